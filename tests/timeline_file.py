"""Reader of the file the library writes when FC_TIMELINE is set: one "name start_us end_us" line per timed kernel or
copy, a "# n spans" line before each collection (used by the FC_TIMELINE test)."""


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
