"""Reader for the small text fixtures under tests/golden/."""
import os

import numpy as np

from paper_2310_09443_amd.traces import Trace

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


class Golden:
    def __init__(self, name):
        self.K = None
        dur, tensors, uses = [], {}, []
        self.params, self.expect = {}, {}
        with open(os.path.join(HERE, name)) as f:
            for line in f:
                line = line.split("#", 1)[0].split()
                if not line:
                    continue
                key, rest = line[0], line[1:]
                if key == "K":
                    self.K = int(rest[0])
                elif key == "dur":
                    dur = [int(x) for x in rest]
                elif key == "tensor":
                    tensors[int(rest[0])] = (int(rest[1]), int(rest[2]))
                elif key == "use":
                    uses.append((int(rest[0]), int(rest[1])))
                elif key == "param":
                    v = [int(x) for x in rest[1:]]
                    self.params[rest[0]] = v if len(v) > 1 else v[0]
                elif key == "expect":
                    self.expect.setdefault(rest[0], []).append([int(x) for x in rest[1:]])
                else:
                    raise ValueError(f"{name}: unknown key {key}")
        assert len(dur) == self.K and sorted(tensors) == list(range(len(tensors)))
        self.trace = Trace(name,
                           np.array(dur, np.uint64),
                           np.array([tensors[i][0] for i in range(len(tensors))], np.uint64),
                           np.array([tensors[i][1] for i in range(len(tensors))], np.uint8),
                           np.array([u[0] for u in uses], np.uint32),
                           np.array([u[1] for u in uses], np.uint32))

    def plan_args(self):
        p = self.params
        return dict(gpu_cap=p["gpu_cap"], host_cap=p["host_cap"], bw_out=p["bw_out"], bw_in=p["bw_in"])

    def variant_args(self):
        """Ranking key and benefit reading of the example (0 / absent: the default)."""
        return dict(rank=self.params.get("rank", 0), area=self.params.get("area", 0))
