"""The PASTA-LANG interpreter's control flow on a synthetic trace -- TEST INFRASTRUCTURE.

What is followed (arxiv 2502.11517, Section 3, "Interpreter" and "Efficiency"; Figure 2): the
interpreter decodes the main thread until a promise tag, starts a thread for it at once (the
inserted <async> token opens the thread's context), keeps decoding all live threads in the same
forward passes, holds a sync token back until the threads have ended, then lets the main thread
go on with everything in its context.  Position ids after a promise are ESTIMATED from the
length the promise predicts (Section 4, "Training a PASTA-SFT model"; appendix "Positional
Embedding").  Written as a little simulation of thread objects, pass by pass; it shares no code
with the library's replay.

Conventions where the paper is silent (same as the library's header): rows of a pass enter the
pool in the order main thread, thread born in this pass, older threads by age; a thread's
</async> token is fed like any other token; a fork takes the lowest free thread id >= 1, ids
become free when the sync that joins them is executed.
"""
from __future__ import annotations

TEXT, PROMISE, SYNC = 0, 1, 2


class _Thread:
    def __init__(self, tid, pos, todo):
        self.tid, self.pos, self.todo = tid, pos, todo  # todo: tokens it still has to feed


def interpret(ops, first_pos, first_slot, max_threads):
    """Returns (tokens, n_passes): tokens in feeding order, each a dict
    {slot, stream, parent, new, join, pos, pass_}; `new` marks a thread's first token (the main
    thread's context, stream 0, exists already: none of its tokens is `new`)."""
    script = []  # the main thread's tokens, one entry each
    for kind, a, b in ops:
        if kind == TEXT:
            script += [("text",)] * a
        elif kind == PROMISE:
            script.append(("promise", a, b))
        else:
            script.append(("sync",))
    tokens, forks, unjoined = [], [], []
    free = list(range(1, max_threads))
    main_pos, i, passes, slot = first_pos, 0, 0, first_slot

    def feed(stream, parent, new, join, pos):
        nonlocal slot
        tokens.append(dict(slot=slot, stream=stream, parent=parent, new=new, join=join, pos=pos, pass_=passes))
        slot += 1

    while i < len(script) or any(f.todo for f in forks):
        older = [f for f in forks if f.todo]
        if i < len(script):
            item = script[i]
            if item[0] == "text":
                feed(0, -1, False, [], main_pos)
                main_pos += 1
                i += 1
            elif item[0] == "promise":
                if not free:
                    raise OverflowError("more threads than ids")
                tid = free.pop(0)
                feed(0, -1, False, [], main_pos)            # the promise
                feed(tid, 0, True, [], main_pos + 1)        # the inserted <async>
                forks.append(_Thread(tid, main_pos + 2, item[2] + 1))
                unjoined.append(tid)
                main_pos += 1 + item[1]                     # estimated ids: skip the predicted length
                i += 1
            elif not older:                                 # sync, and nobody left to wait for
                feed(0, -1, False, list(unjoined), main_pos)
                main_pos += 1
                free = sorted(free + unjoined)
                unjoined, forks = [], []
                i += 1
        for f in older:
            feed(f.tid, -1, False, [], f.pos)
            f.pos += 1
            f.todo -= 1
        passes += 1
    return tokens, passes
