"""Reader of the hand-typed fixture format under tests/golden/ (plain text, no arithmetic)."""
import os

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_fixture(name):
    size = json_text = body = None
    expect, meta, scalars, parts = [], {}, {}, []
    with open(os.path.join(GOLDEN, name), encoding="utf-8") as f:
        for line in f:
            line = line.rstrip("\n")
            if line.startswith("#") or not line.strip():
                continue
            key, _, val = line.partition(": ")
            if key == "size_le":
                size = bytes.fromhex(val.replace(" ", ""))
            elif key == "json":
                json_text = val.encode("utf-8")
            elif key == "body":
                body = bytes.fromhex(val.replace(" ", ""))
            elif key == "expect":
                nm, dt, shape, b, e, hexbytes = val.split(" ")
                shp = () if shape == "-" else tuple(int(x) for x in shape.split(","))
                data = b"" if hexbytes == "-" else bytes.fromhex(hexbytes)
                expect.append((nm, dt, shp, int(b), int(e), data))
            elif key == "expect_part":
                nm, dst, dim, blocks, rank, world, shape, hexbytes = val.split(" ")
                parts.append((nm, None if dst == "-" else dst, int(dim), int(blocks), int(rank), int(world),
                              tuple(int(x) for x in shape.split(",")), bytes.fromhex(hexbytes)))
            elif key == "expect_meta":
                k, v = val.split(" ")
                meta[k] = v
            elif key.startswith("expect_"):
                scalars[key[7:]] = int(val)
    return dict(file=size + json_text + body, expect=expect, meta=meta, parts=parts, **scalars)
