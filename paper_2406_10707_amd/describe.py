"""python -m paper_2406_10707_amd.describe <checkpoint file or directory>: prints the tensor table the
file carries (for a directory: of its newest whole checkpoint). No GPU needed."""
import os
import sys

from . import binding as B


def main(argv):
    if len(argv) != 2:
        print(__doc__)
        return 2
    path = argv[1]
    if os.path.isdir(path):
        _, path = B.find_latest(path)
    sys.stdout.write(path + "\n" + B.describe_file(path))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
