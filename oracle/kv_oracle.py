"""TEST INFRASTRUCTURE -- plain Python statement of the KV page pool with prefix caching.

Only tests/ (and the bench scripts' baseline legs) may import this module; the library never does.

Passages of arxiv 2504.14775 this follows: the KV cache is handed out in pages before a micro-batch runs and all
pipeline stages share one set of page tables (section 3.1, caption of the prefill case study; section 3.3, the
driver worker manages the KV cache); the runtime integrates PagedAttention and prefix caching (section 3.4;
section 5 names the radix-tree reuse of KV across requests as the prior work this comes from).  The paper gives
no algorithm for either, so what follows is a reading, stated once here:

  K1  A page holds 16 tokens.  Only a page that is completely filled with prompt tokens can be shared; it is
      identified by its 16 token ids together with the identity of the page that holds the 16 tokens before
      them (none for the first page): a radix tree over whole pages, so two prompts share exactly their
      longest common prefix of whole pages.  No hashing: two different prefixes can never be confused.
  K2  Every page has a count of the requests that hold it.  A registered page whose count is zero keeps its
      content and waits in an eviction queue; it counts as idle KV memory (it can be reclaimed at once).
  K3  A new page is taken from the free stack (last in, first out; 0, 1, 2, ... at the start) and, when that
      is empty, from the front of the eviction queue: least recently released first, and of the pages one
      request releases together the one deepest in the tree first -- so a page is never evicted before a
      page that extends it.
  K4  A request releases all its pages at once: unregistered pages whose count drops to zero go onto the free
      stack in block-table order, registered ones to the back of the eviction queue, last table entry first.
  K5  A lookup walks the tree along the prompt, takes a count on every page it finds and stops at the first
      page that is missing; the caller bounds the walk so that at least one prompt token is left to compute.
  K6  Registering a page whose key is already present (another request computed the same prefix meanwhile)
      fails and leaves the page private.
"""
from collections import OrderedDict
from typing import List, Optional, Sequence, Tuple

PAGE = 16
ROOT = -1


class PagePool:
    def __init__(self, total_pages: int):
        assert total_pages >= 1
        self.total = total_pages
        self.free: List[int] = list(range(total_pages - 1, -1, -1))        # K3: the top is the end of the list
        self.count = [0] * total_pages
        self.key: List[Optional[Tuple[int, Tuple[int, ...]]]] = [None] * total_pages   # of a registered page
        self.index = {}                                                     # key -> page
        self.children = [0] * total_pages
        self.queue: "OrderedDict[int, None]" = OrderedDict()               # K2: oldest first
        self.evictions = 0

    def available(self) -> int:
        """Pages that alloc() can still hand out: free ones and registered ones nobody holds."""
        return len(self.free) + len(self.queue)

    def alloc(self) -> int:
        assert self.available() > 0
        if self.free:
            page = self.free.pop()
        else:
            page, _ = self.queue.popitem(last=False)
            assert self.children[page] == 0                                 # K3: a leaf of the tree
            parent = self.key[page][0]
            del self.index[self.key[page]]
            self.key[page] = None
            if parent != ROOT:
                self.children[parent] -= 1
            self.evictions += 1
        assert self.count[page] == 0
        self.count[page] = 1
        return page

    def match(self, tokens: Sequence[int], max_pages: int) -> List[int]:
        """K5.  tokens: the prompt; at most max_pages pages are looked up."""
        found: List[int] = []
        parent = ROOT
        for i in range(min(max_pages, len(tokens) // PAGE)):
            page = self.index.get((parent, tuple(tokens[i * PAGE:(i + 1) * PAGE])))
            if page is None:
                break
            found.append(page)
            parent = page
        for page in found:
            if self.count[page] == 0:
                del self.queue[page]
            self.count[page] += 1
        return found

    def register(self, parent: int, tokens16: Sequence[int], page: int) -> bool:
        """K1, K6.  parent: the registered page holding the 16 tokens before these (ROOT for the first page)."""
        assert len(tokens16) == PAGE and self.count[page] >= 1 and self.key[page] is None
        assert parent == ROOT or (self.key[parent] is not None and self.count[parent] >= 1)
        k = (parent, tuple(tokens16))
        if k in self.index:
            return False
        self.index[k] = page
        self.key[page] = k
        if parent != ROOT:
            self.children[parent] += 1
        return True

    def release(self, pages: Sequence[int]) -> None:
        """K4.  pages: a request's block table."""
        for page in pages:
            assert self.count[page] >= 1
            self.count[page] -= 1
            if self.count[page] == 0 and self.key[page] is None:
                self.free.append(page)
        for page in reversed(pages):
            if self.count[page] == 0 and self.key[page] is not None:
                self.queue[page] = None
