"""Writes closed_forms.txt: values that Eq. (1) and the image-method definition fix in closed form.

The paper prints no worked numerical example for this path, so the fixtures are special cases that can
be evaluated by hand.  Only Python's math module is used here: nothing from oracle/ or from the library.

  warp  alpha  omega  omega'     Eq. (1) at omega = 0, pi/2, pi, where sin and cos are 0 or +-1:
                                 omega'(0) = 0, omega'(pi) = pi, omega'(pi/2) = pi/2 + 2 atan(1 - alpha);
                                 and at omega = pi/3 (sin = sqrt(3)/2, cos = 1/2).
  direct  r  fs  c  tap  amplitude   beta = 0 leaves the direct path only (Sec. 2.3's simulator):
                                 one impulse 1 / (4 pi r) at tap floor(r fs / c + 1/2).
  mel  f_hz  mel                 2595 log10(1 + f / 700) at f = 0, 700, 6300 (log10 of 1, 2, 10).
"""
import math
import os


def main():
    lines = ["# kind, then the columns named in make_closed_forms.py"]
    for alpha in (0.8, 0.9, 1.0, 1.1, 1.2):
        a = 1.0 - alpha
        lines.append(f"warp {alpha!r} 0.0 0.0")
        lines.append(f"warp {alpha!r} {math.pi / 2!r} {math.pi / 2 + 2.0 * math.atan(a)!r}")
        lines.append(f"warp {alpha!r} {math.pi!r} {math.pi!r}")
        w = math.pi / 3
        lines.append(f"warp {alpha!r} {w!r} {w + 2.0 * math.atan(a * math.sqrt(3.0) / 2.0 / (1.0 - a / 2.0))!r}")
    for r, fs, c in ((1.0, 16000.0, 343.0), (2.5, 16000.0, 343.0), (7.25, 16000.0, 340.0), (0.3, 8000.0, 343.0)):
        lines.append(f"direct {r!r} {fs!r} {c!r} {math.floor(r * fs / c + 0.5)} {1.0 / (4.0 * math.pi * r)!r}")
    for f, m in ((0.0, 0.0), (700.0, 2595.0 * math.log10(2.0)), (6300.0, 2595.0)):
        lines.append(f"mel {f!r} {m!r}")
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "closed_forms.txt"), "w") as fh:
        fh.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
