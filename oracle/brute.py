"""Pure-Python brute force of the 3x3x3 'same' convolution (test infrastructure only).

Independent of the C oracle and deliberately written the other way round: in
scatter form.  Every input voxel pushes its contribution through every tap to the
output voxel that would read it, one multiply-add at a time on nested lists.  A
sign or index slip in the gather-form C loops does not survive the comparison.
"""


def conv3d_same_scatter(x, w, bias=None):
    """x[N][D][H][W][Cin], w[3][3][3][Cin][Cout] as nested lists -> y nested lists."""
    N, D, H, W, Cin = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0]), len(x[0][0][0][0])
    Cout = len(w[0][0][0][0])
    y = [[[[[(0.0 if bias is None else bias[co]) for co in range(Cout)] for _ in range(W)]
           for _ in range(H)] for _ in range(D)] for _ in range(N)]
    for n in range(N):
        for sd in range(D):
            for sh in range(H):
                for sw in range(W):
                    for kd in range(3):
                        for kh in range(3):
                            for kw in range(3):
                                # the output voxel whose tap (kd,kh,kw) lands on (sd,sh,sw)
                                d, h, ww = sd - (kd - 1), sh - (kh - 1), sw - (kw - 1)
                                if not (0 <= d < D and 0 <= h < H and 0 <= ww < W):
                                    continue
                                for ci in range(Cin):
                                    xv = x[n][sd][sh][sw][ci]
                                    for co in range(Cout):
                                        y[n][d][h][ww][co] += xv * w[kd][kh][kw][ci][co]
    return y
