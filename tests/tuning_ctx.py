"""Context manager for the library's process-wide tuning keys (usable without a GPU)."""
import paper_2410_22249_amd as emb


class tuning:
    """Set tuning keys, restore the previous values on exit."""

    def __init__(self, **kw):
        self.kw = kw
        self.old = {}

    def __enter__(self):
        for k, v in self.kw.items():
            self.old[k] = emb.emb_bag_get_tuning(k)
            emb.emb_bag_set_tuning(k, v)
        return self

    def __exit__(self, *exc):
        for k, v in self.old.items():
            emb.emb_bag_set_tuning(k, v)
        return False
