"""Reads the file the library writes when FC_TIMELINE is set (one "name start_us end_us" line per timed kernel or copy,
a "# n spans" line before each collection) and prints, for the first collection, the spacing of the miss-fill launches
and every span of a window of three fetches in start order.

    FC_TIMELINE=/tmp/tl.txt python bench.py --profile-steps 20 --cpu-batches 0
    python -m paper_2208_05321_amd.timeline /tmp/tl.txt [index of the first fetch of the window]
"""
import sys


def load_first_collection(path):
    spans, seen = [], 0
    with open(path) as f:
        for line in f:
            if line.startswith("#"):
                seen += 1
                if seen > 1:
                    break
                continue
            name, a, b = line.split()
            spans.append((float(a), float(b), name))
    spans.sort()
    return spans


def main(argv):
    spans = load_first_collection(argv[1])
    first = int(argv[2]) if len(argv) > 2 else 10
    fills = [s for s in spans if s[2] == "miss_fill"]
    print(f"{len(spans)} spans, {len(fills)} miss fills")
    for i in range(max(1, first - 2), min(len(fills), first + 6)):
        a, b, _ = fills[i]
        pb = fills[i - 1][1]
        print(f"fill {i}: start {a:.0f} us, lasts {b - a:.0f}, idle before it {a - pb:.0f}, end to end {b - pb:.0f}")
    if first + 2 >= len(fills):
        return
    t0, t1 = fills[first][0], fills[first + 2][1]
    print(f"\nstart / end / duration (us, relative to the start of fill {first}):")
    for a, b, name in spans:
        if t0 - 50 <= a <= t1:
            print(f"{a - t0:8.0f} {b - t0:8.0f} {b - a:7.0f}  {name}")


if __name__ == "__main__":
    main(sys.argv)
