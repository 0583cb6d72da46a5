"""Lines that the tests want in the run's summary (what was covered, how long it took), shown
at the end of the session also when output capture hides the tests' own prints."""
LINES = []


def note(msg: str) -> None:
    LINES.append(msg)
    print(msg, flush=True)
