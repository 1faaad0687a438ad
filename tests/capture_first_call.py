"""Run as a program in a fresh process (test_gpu_launch_modes.py starts it): the first stage calls this process ever
makes - the draft module's layer, the draft head, collapse/tree, the Eq. 5 values, verification attention, the base
head, acceptance and the history update - are recorded by a stream capture right after ctcspec_create, replayed, and
compared bit for bit with eager calls made afterwards."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)
sys.path.insert(0, os.path.dirname(HERE))


def main():
    import paper_2412_00061_amd as pkg
    pkg.load_library()
    from test_gpu_launch_modes import whole_decode_step_graph_replay
    whole_decode_step_graph_replay(pkg, capture_first=True)
    print("capture-first ok", flush=True)


if __name__ == "__main__":
    main()
