#!/usr/bin/env python3
"""Writes the two derived fixtures of this folder from the numbers the paper prints.

    python tests/golden/make_fixtures.py          # rewrite the files
    python tests/golden/make_fixtures.py --check  # exit 1 if a committed file differs

Nothing here calls the library or the oracle: every stored value is either printed in the paper
(arxiv 2502.11517, Section 3, paragraph "Efficiency", the walk through Figure 2: pool indices
i = 19-20 at T=0 and i = 26-27 at T=3; Fork#2 ends at T=22, Fork#1 at T=34; then the sync token
enters the pool) or follows from those by the counting written out below.

paper_sec3_sync.json  continues paper_sec3_visibility.json (one pool slot per token; inside T=2 the
order Fork#1 token, second promise, second <async>) up to the sync token:
  slots 0..27   as in paper_sec3_visibility.json;
  T=3..22       both forks decode: T=k puts Fork#1's token in slot 26 + 2 (k - 3) and Fork#2's in the
                next slot (the printed pair i = 26-27 is k = 3), so Fork#2's last token (T=22) is slot 65;
  T=23..34      Fork#1 alone: slots 66..77;
  slot 78       the sync token of the main thread, joining both forks.
The facts are slots picked by hand whose visibility the text states: after the sync the main thread
sees everything; before it no thread sees another thread's tokens, a fork sees the main thread's
tokens up to its own spawn (Fork#2 therefore both promises, Fork#1 only the first).

paper_sec3_replay.json  the same timeline as a trace (promise, promise, sync, three text tokens) under
the feeding order of the replay (main thread, thread born in this pass, older threads by age).  A
fork born in pass p feeds its <async> token in pass p and its b content tokens plus </async> in the
b + 1 passes after it, so content lengths 32 and 19 end Fork#1 in pass 33 and Fork#2 in pass 21
(the text's T=34 and T=22, passes counted from 0).
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))

N_PROMPT = 21            # slots 0..20: the text's i = 19-20 are the prompt's last two
T_PAIR, SLOT_PAIR = 3, 26  # "i = 26-27" at T=3
T_FORK2_END, T_FORK1_END = 22, 34


def sync_fixture():
    vis = json.load(open(os.path.join(HERE, "paper_sec3_visibility.json")))
    ev_stream = list(vis["slot_stream"])                    # slots 0..27
    assert len(ev_stream) == SLOT_PAIR + 2
    ev_parent = [-1] * len(ev_stream)
    ev_new = [0] * len(ev_stream)
    ev_new[0] = 1
    for sid, name in ((1, "fork1"), (2, "fork2")):          # a thread's first slot carries its parent
        first = ev_stream.index(sid)
        ev_parent[first], ev_new[first] = vis["stream_parent"][sid], 1
    for T in range(T_PAIR + 1, T_FORK2_END + 1):            # both forks, alternating
        ev_stream += [1, 2]
    for T in range(T_FORK2_END + 1, T_FORK1_END + 1):       # Fork#1 alone
        ev_stream += [1]
    sync_slot = len(ev_stream)
    ev_stream += [0]
    ev_parent += [-1] * (len(ev_stream) - len(ev_parent))
    ev_new += [0] * (len(ev_stream) - len(ev_new))
    f2_last = SLOT_PAIR + 2 * (T_FORK2_END - T_PAIR) + 1
    assert ev_stream[f2_last] == 2 and 2 not in ev_stream[f2_last + 1:]
    f1_last = sync_slot - 1
    return {
        "citation": "arxiv 2502.11517, Section 3, paragraph 'Efficiency': the two forks alternate in the pool from T=3 to "
                    "T=22, Fork#2 ends at T=22 and Fork#1 at T=34, then the <sync/> token enters the pool and the main "
                    "thread resumes 'conditioning on both forks' asynchronous generations'; the attention-mask paragraph: "
                    "a token attends to any ancestor reachable backwards along Figure 2b's edges, and threads cannot "
                    "attend to each other's tokens before synchronization.",
        "assumption": "continues tests/golden/paper_sec3_visibility.json (one slot per token).  With this count the "
                      "<sync/> token lands in slot 78; the text prints i=80 (the figure that would settle the two missing "
                      "slots is not in the text), so only the STRUCTURE is used: who sees what.",
        "ev_stream": ev_stream, "ev_parent": ev_parent, "ev_new": ev_new,
        "join": {str(sync_slot): [1, 2]},
        "sync_slot": sync_slot,
        "facts": [
            {"query_slot": sync_slot, "sees_all_slots_up_to_itself": True},
            {"query_slot": f1_last,
             "note": "Fork#1's last token: prompt, first promise, its own tokens; nothing of Fork#2, not the second promise",
             "must_see": [0, 20, 21, 22, 23, 26, 28, f2_last + 1, f1_last],
             "must_not_see": [24, 25, 27, 29, f2_last]},
            {"query_slot": f2_last,
             "note": "Fork#2's last token (T=22): sees both promises, none of Fork#1",
             "must_see": [21, 24, 25, 27, 29, f2_last - 2],
             "must_not_see": [22, 23, 26, 28, f2_last - 1]},
        ],
    }


def replay_fixture():
    # content tokens so that the forks end where the text says (a fork born in pass p ends in pass p + b + 1)
    b1 = (T_FORK1_END - 1) - 0 - 1
    b2 = (T_FORK2_END - 1) - 1 - 1
    ops = [[1, 30, b1], [1, 20, b2], [2, 0, 0], [0, 3, 0]]  # predicted lengths: multiples of ten near the real ones
    n_text = 3
    n_tokens = n_text + 1 + (3 + b1) + (3 + b2)             # text, sync, per promise: promise + <async> + b + </async>
    sync_pass = (T_FORK1_END - 1) + 1                        # the pass after the last fork's last
    return {
        "citation": "arxiv 2502.11517, Section 3, paragraph 'Efficiency' (the walk through Figure 2): promise at T=1 with "
                    "the interpreter-inserted <async> right behind it; at T=2 Fork#1 decodes while a second promise starts "
                    "Fork#2; at T=3 three tokens are decoded in parallel from three threads, of which the <sync/> token "
                    "does not enter the pool until later while the other two enter at neighbouring positions i=26-27; the "
                    "forks alternate until Fork#2 ends at T=22 and Fork#1 at T=34; then the <sync/> token enters the pool "
                    "and the main thread resumes conditioning on both forks.",
        "assumption": "prompt in slots 0-20 (the text's i=19-20 are its last two); a token decoded at timestamp T is fed, "
                      "and enters the pool, in the following pass.  With this count the <sync/> token lands in slot 78; "
                      "the text prints i=80 (the figure that would settle it is not in the text): only the structure is "
                      "pinned.",
        "n_prompt": N_PROMPT,
        "ops": ops,
        "facts": {
            "pass0_slots": {"21": "promise #1 (main)", "22": "<async> #1 (Fork#1)"},
            "pass0": [[21, 0], [22, 1]],
            "pass1": [[23, 0], [24, 2], [25, 1]],
            "pass2": [[SLOT_PAIR, 1], [SLOT_PAIR + 1, 2]],
            "three_threads_decode_in_pass1": True,
            "fork2_last_pass": T_FORK2_END - 1, "fork1_last_pass": T_FORK1_END - 1,
            "sync_slot": N_PROMPT + n_tokens - 1 - n_text, "sync_pass": sync_pass, "sync_joins": [1, 2],
            "n_tokens": n_tokens, "n_passes": sync_pass + 1 + n_text,
        },
    }


def main():
    check = "--check" in sys.argv[1:]
    bad = 0
    for name, obj, indent in (("paper_sec3_sync.json", sync_fixture(), 1), ("paper_sec3_replay.json", replay_fixture(), 1)):
        path = os.path.join(HERE, name)
        if check:
            same = json.load(open(path)) == obj
            print(name, "matches" if same else "DIFFERS")
            bad += not same
        else:
            with open(path, "w") as f:
                json.dump(obj, f, indent=indent)
                f.write("\n")
            print("wrote", path)
    sys.exit(1 if bad else 0)


if __name__ == "__main__":
    main()
