"""The token rules of the CML stream (Sec. 3 and Sec. 5.1), written for the tests as a function of the whole generated
history instead of an incremental state machine: the oracle replays of the end-to-end session tests use this and not
the product's monitor, and a host test checks the two against each other on random streams.

A call block is  CALL id.. HEAD body.. END,  a trap  TRAP END;  interrupt blocks are never generated (they are
appended by the interrupt manager and are not part of this history).
"""


def _where(generated, cml):
    """('text' | 'id' | 'body' | 'trap', id tokens, body tokens) after the generated tokens."""
    where, ids, body = "text", [], []
    for t in generated:
        if where == "text":
            if t == cml.call:
                where, ids, body = "id", [], []
            elif t == cml.trap:
                where = "trap"
        elif where == "id":
            if t == cml.head:
                where = "body"
            else:
                ids.append(t)
        elif where == "body":
            if t == cml.end:
                where = "text"
            else:
                body.append(t)
        else:                       # the END that closes a trap
            where = "text"
    return where, ids, body


class ReferenceMonitor:
    def __init__(self, cml):
        self.cml = cml
        self.generated = []

    @property
    def critical(self):
        """Inside a block no interrupt may be inserted (Sec. 3.2)."""
        return _where(self.generated, self.cml)[0] != "text"

    def banned(self):
        c, where = self.cml, _where(self.generated, self.cml)[0]
        return {"text": [c.intr, c.head, c.end],           # only CALL or TRAP open a block; INTR is never generated
                "id": [c.call, c.intr, c.trap, c.end],     # an identifier ends with HEAD
                "body": [c.call, c.intr, c.trap, c.head],  # a body ends with END
                "trap": [c.intr]}[where]

    def forced(self):
        return self.cml.end if _where(self.generated, self.cml)[0] == "trap" else None

    def observe(self, token):
        before, ids, body = _where(self.generated, self.cml)
        self.generated.append(int(token))
        after = _where(self.generated, self.cml)[0]
        if before == "body" and after == "text":
            return ("call", ids, body)
        if before == "trap":
            return ("trap",)
        return None
