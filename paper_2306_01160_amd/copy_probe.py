"""Plain copy of known size, for calibrating rocprofv3's FETCH_SIZE / WRITE_SIZE counters.

    python -m paper_2306_01160_amd.copy_probe [S T d]

Runs scfa_gather_rows with the identity index (out[s,r,:] = x[s,r,:], same dtype): per launch it
reads S*T*(2d + 4) bytes and writes S*T*2d bytes.  Prints those two figures.
"""
import sys

import torch

from . import binding as sc


def main():
    S, T, d = (int(a) for a in sys.argv[1:4]) if len(sys.argv) >= 4 else (24, 16384, 64)
    dev = torch.device("cuda:0")
    x = torch.randn((S, T, d), device=dev).to(torch.bfloat16)
    idx = torch.arange(T, dtype=torch.int32, device=dev).repeat(S, 1).contiguous()
    out = torch.empty_like(x)
    for _ in range(10):
        sc.scfa_gather_rows(x, idx, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out, x)
    print(f"copy_probe: per launch reads {S * T * (2 * d + 4)} bytes, writes {S * T * 2 * d} bytes")


if __name__ == "__main__":
    main()
