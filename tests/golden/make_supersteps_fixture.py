#!/usr/bin/env python3
"""Writes ``worked_examples_supersteps.json`` next to this file.

The inputs below were chosen, and their ``by_hand`` notes worked out, on paper for this library's reading of a run of
supersteps (Fig. 1 and Section III of the ElasticBSP paper describe it in words only).  The expected barriers, waits and
iteration counts stored in the fixture are computed here by ``oracle.simulate`` and by nothing else: no GPU code is
imported.  ``tests/test_oracle_simulate.py`` checks that the committed fixture is what this script writes.

    python tests/golden/make_supersteps_fixture.py
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

SOURCE = ("inputs and by_hand notes worked on paper for this library's reading of a run of supersteps (Fig. 1 and Section III "
          "of the ElasticBSP paper describe it in words only); expected values computed by oracle.simulate in "
          "tests/golden/make_supersteps_fixture.py")

CASES = [
    {
        "name": "two workers, iteration times 2 and 3, R = 3: they meet at 6 without waiting, again and again",
        "last_end0": [
            [
                0,
                0
            ]
        ],
        "interval": [
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    2,
                    3
                ]
            ]
        ],
        "R": 3,
        "sync_cost": 0,
        "by_hand": "rows (2,4,6) and (3,6,9); candidates >= 3: c=3 -> (3-2)+0 = 1, c=4 -> 0+(4-3) = 1, c=6 -> 0, c=9 -> (9-6)+0 = 3"
    },
    {
        "name": "the same with a synchronisation of 5 after every barrier",
        "last_end0": [
            [
                0,
                0
            ]
        ],
        "interval": [
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    2,
                    3
                ]
            ]
        ],
        "R": 3,
        "sync_cost": 5,
        "by_hand": "every worker restarts at barrier + 5: 6 + 5 = 11, 11 + 6 = 17, 17 + 5 + 6 = 28"
    },
    {
        "name": "R = 2 cannot reach the meeting point: the first minimum is the first candidate",
        "last_end0": [
            [
                0,
                0
            ]
        ],
        "interval": [
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    2,
                    3
                ]
            ]
        ],
        "R": 2,
        "sync_cost": 0,
        "by_hand": "rows (2,4) and (3,6); c=3 -> 1, c=4 -> 1, c=6 -> (6-4)+0 = 2: barrier 3, wait 1"
    },
    {
        "name": "different start times only matter in the first superstep",
        "last_end0": [
            [
                1,
                0
            ]
        ],
        "interval": [
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    2,
                    3
                ]
            ]
        ],
        "R": 3,
        "sync_cost": 0,
        "by_hand": "rows (3,5,7) and (3,6,9): c=3 -> 0; from 3 on the pattern of the first case"
    },
    {
        "name": "iteration times change between supersteps",
        "last_end0": [
            [
                0,
                0
            ]
        ],
        "interval": [
            [
                [
                    2,
                    3
                ]
            ],
            [
                [
                    4,
                    2
                ]
            ]
        ],
        "R": 2,
        "sync_cost": 1,
        "by_hand": "superstep 1 starts at 3 + 1 = 4: rows (8,12) and (6,8); candidates >= 8: c=8 -> 0+0"
    },
    {
        "name": "R = 1 is BSP: the slowest worker sets every barrier",
        "last_end0": [
            [
                0,
                0,
                0
            ]
        ],
        "interval": [
            [
                [
                    5,
                    7,
                    6
                ]
            ],
            [
                [
                    4,
                    4,
                    9
                ]
            ]
        ],
        "R": 1,
        "sync_cost": 2,
        "by_hand": "superstep 0: ends 5,7,6 -> barrier 7, wait 2+0+1; restart at 9: ends 13,13,18 -> barrier 18, wait 5+5+0"
    }
]


def build():
    import oracle
    out = []
    for c in CASES:
        barrier, iters, wait, rc, _ = oracle.simulate(np.array(c["last_end0"], dtype=np.int64), np.array(c["interval"], dtype=np.int64),
                                                      c["R"], c["sync_cost"], threads=1)
        assert (rc == 0).all()
        out.append({"name": c["name"], "last_end0": c["last_end0"], "interval": c["interval"], "R": c["R"], "sync_cost": c["sync_cost"],
                    "barrier": barrier.tolist(), "wait": wait.tolist(), "iters": iters.tolist(), "by_hand": c["by_hand"]})
    return {"source": SOURCE, "cases": out}


if __name__ == "__main__":
    with open(os.path.join(HERE, "worked_examples_supersteps.json"), "w") as f:
        json.dump(build(), f, indent=1)
        f.write("\n")
