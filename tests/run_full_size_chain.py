#!/usr/bin/env python3
"""A configuration's whole chain at full size against the oracle, outside pytest (the oracle's full sort
makes the ResNet-50 and VGG-16 shapes take a quarter of an hour, too long for the GPU suite, which
runs them at a sixteenth of the row length instead).  Every step compares the descriptors, the server
error and every model row bit for bit and stops at the first mismatch.

    python tests/run_full_size_chain.py c4_resnet50_topk [steps]
"""
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main() -> int:
    import test_gpu_fullsize as T

    name = sys.argv[1] if len(sys.argv) > 1 else "c4_resnet50_topk"
    w = T.WL[name]
    steps = int(sys.argv[2]) if len(sys.argv) > 2 else w.steps
    t0 = time.time()
    T._chain(w, steps, f"whole chain, full size {name}", progress_every=1,
             expect_slow_rows=0 if "topk" in (w.worker_comp, w.server_comp) else None)
    print(f"RESULT {name}: {steps} chained steps at N={w.N} d={w.d} bit-identical to the oracle "
          f"({time.time() - t0:.0f} s)", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
