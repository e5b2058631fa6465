"""Times the single-GEMM entry points (ah_gemm_nn / nt / tn) on one shape, for operand data of a
chosen kind.  The MFMA rate of an MI355X is limited by board power, and the power of a matrix
multiplication depends on how many operand bits toggle: the same kernel on the same shape is much
faster on constant or zero data than on random data.  This tool shows both numbers.

Usage (on an MI355X):  python -m paper_2512_20953_amd.gemm_probe --layout nn --shape 4096 8192 4096 --data normal constant zero
With --library the same products are also timed through torch.matmul (the vendor's GEMM library), as a
reference for what a tuned GEMM reaches on this board and data; the library is not part of the stage path.
"""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def time_gemm(layout, M, N, K, data, iters=1000, library=False):
    import torch
    import paper_2512_20953_amd as P

    def make(shape, std):
        if data == "normal":
            return (torch.randn(*shape, device="cuda") * std).to(torch.bfloat16)
        if data == "constant":
            return torch.full(shape, std, device="cuda", dtype=torch.bfloat16)
        return torch.zeros(*shape, device="cuda", dtype=torch.bfloat16)

    if layout == "nn":
        A, B, C = make((M, K), 1.0), make((K, N), 0.02), torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
        run = lambda: P.gemm_nn(A, B, None, C)
    elif layout == "nt":
        A, B, C = make((M, K), 1.0), make((N, K), 0.02), torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
        run = lambda: P.gemm_nt(A, B, C)
    else:
        A, B, C = make((K, M), 1.0), make((K, N), 1.0), torch.zeros(M, N, device="cuda", dtype=torch.float32)
        run = lambda: P.gemm_tn(A, B, C, 1)
    if library:
        if layout == "nn":
            run = lambda: torch.matmul(A, B, out=C)
        elif layout == "nt":
            run = lambda: torch.matmul(A, B.t(), out=C)
        else:
            Cb = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)   # bf16 output: the library has no fp32 accumulate-in-place
            run = lambda: torch.matmul(A.t(), B, out=Cb)
    for _ in range(20):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    return ms * 1e3, 2.0 * M * N * K / (ms * 1e-3) / 1e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layout", nargs="+", default=["nn", "nt", "tn"])
    ap.add_argument("--shape", type=int, nargs=3, default=[4096, 8192, 4096], metavar=("M", "N", "K"))
    ap.add_argument("--data", nargs="+", default=["normal", "constant", "zero"])
    ap.add_argument("--iters", type=int, default=1000)
    ap.add_argument("--library", action="store_true", help="also time torch.matmul on the same operands")
    args = ap.parse_args()
    M, N, K = args.shape
    print("| kernel | layout | M | N | K | operand data | us per launch | TFLOP/s | % of 2500 |")
    print("|---|---|---|---|---|---|---|---|---|")
    for lay in args.layout:
        for d in args.data:
            for lib in ([False, True] if args.library else [False]):
                us, tf = time_gemm(lay, M, N, K, d, args.iters, lib)
                print("| %s | %s | %d | %d | %d | %s | %.1f | %.0f | %.1f |" % ("torch.matmul" if lib else "ah_gemm", lay, M, N, K, d, us, tf, tf / 25.0),
                      flush=True)


if __name__ == "__main__":
    main()
