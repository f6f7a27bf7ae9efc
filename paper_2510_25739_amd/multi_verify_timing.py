"""Times hawk_multi_verify on synthetic logit rows (the figures quoted in the design notes and the
profile summary): python -m paper_2510_25739_amd.multi_verify_timing [config]"""
import json
import sys


def main():
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    import synth
    import paper_2510_25739_amd as H
    s = synth.CONFIGS[int(sys.argv[1]) if len(sys.argv) > 1 else 2]
    out = {"m2": bench.bench_multi_verify(H, s, rows_list=(1, 6, 32, 192), m=2),
           "m4": bench.bench_multi_verify(H, s, rows_list=(6, 192), m=4)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
